"""MI355X-native working-memory decoding path (prune plan, KV compaction with
RoPE re-rotation, paged GQA decode attention) behind a C-ABI library.

`paper_2507_16784_amd.tim` binds the library; importing it fails loudly when
the HIP library has not been built.  `paper_2507_16784_amd.workload` holds the
seeded input generators."""
