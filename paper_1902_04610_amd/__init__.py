"""MI355X-native packed-iteration and job-switch path for Salus-style GPU sharing.

Importing the package is cheap and loads nothing; ``paper_1902_04610_amd.salus``
is the binding of the C-ABI library, ``paper_1902_04610_amd.synth`` the seeded
input generators.
"""
