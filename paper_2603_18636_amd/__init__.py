"""MI355X-native online stage of SVOO (block-sparse 3-D attention for video DiTs).

``paper_2603_18636_amd.svoo`` is the thin binding over the C-ABI library ``libsvoo.so`` (built
from ``csrc/`` by ``build.py``); ``paper_2603_18636_amd.synth`` draws the seeded synthetic inputs.
Importing the package loads nothing native; the binding raises if the library is missing.
"""
