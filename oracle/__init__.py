"""TEST INFRASTRUCTURE: slow, plain CPU oracle for the planner and the stage.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
package.  It shares no code with the product package and never imports it.
"""
