"""TAGC oracle: plain CPU implementation used only to check the HIP library.
Test infrastructure -- never imported by the product package."""
