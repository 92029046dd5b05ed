"""CPU oracle for the RaggedShard / DBuffer hot path.

TEST INFRASTRUCTURE ONLY.  Plain, slow, obviously-correct numpy / pure-Python
definitions of what the path computes (layout plan, ragged_pack, shard_reduce,
FP8 block_quant, dequant_unpack), written from the paper's Section 4 (RaggedShard),
Section 5 (problem statement, Algorithm 1, DBuffer) and the FP8 E4M3 format definition.

Nothing in the product package imports this; it shares no code, tables or constants
with the HIP library.  Only tests, the smoke check and the bench's cpu_baseline leg
may call it.
"""
