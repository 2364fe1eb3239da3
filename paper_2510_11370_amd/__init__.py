"""MI355X-native hot path of Rollout Routing Replay (arxiv 2510.11370, Section 4.1).

``r3``    - thin binding over the C-ABI library (HIP kernels for gfx950).
``synth`` - seeded synthetic inputs (no method arithmetic).
"""
