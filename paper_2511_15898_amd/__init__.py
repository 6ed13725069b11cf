"""MI355X-native Global Resolution verifier (hand-written HIP behind a C ABI).

Importing the package loads nothing; `paper_2511_15898_amd.binding` loads the built library on
first use and fails loudly if it is missing."""
