"""MI355X-native evaluator for batches of candidate request-to-replica assignments.

``binding`` mirrors the C ABI of ``include/autopoiesis_eval.h``; ``traces`` draws the
seeded synthetic inputs; ``build`` compiles the HIP library in-tree.
"""
