"""Batched allocator trace replay on MI355X (GMLake's virtual memory stitching vs. the
splitting caching allocator).  `binding` wraps the C ABI of libvmsreplay.so; `tracegen`
makes the seeded synthetic traces.  Nothing is imported eagerly."""
