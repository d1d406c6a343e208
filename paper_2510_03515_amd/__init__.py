"""MI355X-native fused importance-weighted group-advantage policy-gradient loss (RAPID,
arXiv 2510.03515): thin Python binding over the C-ABI library built from csrc/.

Importing the package does not load the HIP library; `paper_2510_03515_amd.binding` does, on
first use, and raises if it has not been built."""
