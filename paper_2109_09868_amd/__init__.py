"""MI355X-native coding layer of ApproxIFER (arXiv 2109.09868): Berrut encoder,
decoder and Byzantine decoder behind a C ABI.  `paper_2109_09868_amd.binding` loads
the HIP library; `paper_2109_09868_amd.synthetic` draws seeded workloads."""
