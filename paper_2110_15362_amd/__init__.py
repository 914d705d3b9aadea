"""libbittrain: the BitTrain sparse bitmap activation codec for MI355X (gfx950).

``paper_2110_15362_amd.bittrain`` is the thin binding over the C-ABI library
``libbittrain.so`` (hand-written HIP kernels); ``paper_2110_15362_amd.workloads``
draws the seeded synthetic inputs.  Nothing here computes on the CPU: if the
HIP library is missing every call raises.
"""
