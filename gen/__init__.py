"""Seeded synthetic inputs for the JoT finalization pass.

This package only produces inputs (logit rows, initial canvases, planted-token
trajectories).  It contains none of the method's arithmetic (no softmax, no
threshold, no decision) and is the one module both the CPU oracle's tests and
the GPU tests may share.
"""
