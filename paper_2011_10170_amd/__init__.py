"""MI355X-native pattern-sparse 3x3 convolution (forward, backward-data, backward-weight)
with importance-based pattern selection and packing, behind the C-ABI library libpatconv.

Importing the package loads nothing; the binding loads the HIP library on first use and
raises if it is missing (there is no CPU fallback)."""
