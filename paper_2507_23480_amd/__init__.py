"""MI355X-native farthest point sampling, minimum-distance-prediction sampling
and ball query (FastPoint, arXiv 2507.23480).  The HIP library is loaded on
first use by :mod:`paper_2507_23480_amd.binding`; importing this package or
:mod:`paper_2507_23480_amd.inputs` needs no GPU."""
