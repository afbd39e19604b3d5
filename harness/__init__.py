"""Host-side test harness: a reference-counted KV block manager and the seeded
synthetic workload generators that feed both the CPU oracle and the HIP path.

Nothing in this package computes attention or touches cache *contents* beyond
filling them with seeded random numbers: it only produces block tables,
context lengths, slot mappings, copy-on-write pair lists and input values.
"""
