"""MI355X-native batched exact 0/1 multiple-knapsack solver (DeFT's scheduling
core, arXiv 2503.16815).  `workloads` draws synthetic inputs and needs numpy
only; `binding` is the thin wrapper over the C ABI and needs torch + a GPU."""
