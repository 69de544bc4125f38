"""MI355X-native cosine-similarity linear attention (forward and backward).

`binding` wraps the C-ABI library (HIP kernels for gfx950); `autograd` puts
torch.autograd plumbing around it; `inputs` draws the seeded synthetic batches.  Importing this package does not load the library.
"""
